"""The five benchmark workloads: tenant mixes, batch, storage type, input distribution, seed."""
from dataclasses import dataclass
from typing import List, Tuple
from . import zoo


@dataclass
class Config:
    name: str
    dtype: str
    batch: int
    tenants: Tuple[str, ...]
    input_dist: str
    seed: int
    n_stages: int          # stages of the searched schedule

    def models(self):
        return [zoo.BUILDERS[t](self.dtype, self.batch) for t in self.tenants]


CONFIGS = {
    "cfg1": Config("cfg1", "f32", 1, ("tinyA", "tinyB", "tinyC"), "uniform", 101, 2),
    "cfg2": Config("cfg2", "f16", 1, ("resnet18", "vgg16", "mobilenetv2"), "normal", 202, 4),
    "cfg3": Config("cfg3", "f16", 8, ("resnet18", "resnet50", "vgg16", "mobilenetv2"), "normal", 303, 4),
    "cfg4": Config("cfg4", "bf16", 1, ("resnet101", "inceptionv3", "mobilenetv2", "alexnet"), "normal", 404, 4),
    "cfg5": Config("cfg5", "bf16", 16, ("resnet50",) * 8, "normal", 505, 8),
}
