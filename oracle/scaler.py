"""Dynamic loss-scale policy (oracle; test infrastructure only).

Paper Sec. 5 sketches it: raise or lower the factor by watching the weight
gradients for overflow, skipping the update on overflow.  The paper fixes no
constants; the reading used: halve on overflow and reset the clean-step count;
otherwise count the clean step and, once `growth_interval` consecutive clean
steps have been applied, double the factor and reset the count (so the step
after the interval-th clean one already sees the doubled factor).  The factor
is clamped to [min_scale, max_scale].
"""
from dataclasses import dataclass


@dataclass
class Scaler:
    scale: float = 65536.0
    good_steps: int = 0
    growth_interval: int = 1000
    growth: float = 2.0
    backoff: float = 0.5
    min_scale: float = 1.0
    max_scale: float = 16777216.0

    @property
    def inv_scale(self):
        return 1.0 / self.scale

    def update(self, overflow):
        if overflow:
            self.scale = max(self.scale * self.backoff, self.min_scale)
            self.good_steps = 0
        else:
            self.good_steps += 1
            if self.good_steps == self.growth_interval:
                self.scale = min(self.scale * self.growth, self.max_scale)
                self.good_steps = 0
        return self.scale
