"""The five benchmark workloads and the paper's tenant mixes: tenants, batch, storage type, input distribution, seed."""
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


# The tenant combinations of the paper's scalability tables (Tables I-II: two, three and five models, batch 1,
# 224 x 224 inputs), as extra workloads; fp16 storage like cfg2.
PAPER_MIXES = {
    "mix_vgg_r18": Config("mix_vgg_r18", "f16", 1, ("vgg16", "resnet18"), "normal", 611, 4),
    "mix_r18_r34": Config("mix_r18_r34", "f16", 1, ("resnet18", "resnet34"), "normal", 612, 4),
    "mix_r34_r50": Config("mix_r34_r50", "f16", 1, ("resnet34", "resnet50"), "normal", 613, 4),
    "mix_r50_r101": Config("mix_r50_r101", "f16", 1, ("resnet50", "resnet101"), "normal", 614, 4),
    "mix_vgg_r18_r50": Config("mix_vgg_r18_r50", "f16", 1, ("vgg16", "resnet18", "resnet50"), "normal", 615, 4),
    "mix_r18_r34_r50": Config("mix_r18_r34_r50", "f16", 1, ("resnet18", "resnet34", "resnet50"), "normal", 616, 4),
    "mix_5": Config("mix_5", "f16", 1, ("vgg16", "resnet18", "resnet34", "resnet50", "resnet101"), "normal", 617, 4),
}

# Operator-set completion: grouped convolution, local response normalisation and a stand-alone add.
EXTRA = {
    "ops_f32": Config("ops_f32", "f32", 2, ("tinyD", "tinyA"), "uniform", 701, 2),
    "ops_f16": Config("ops_f16", "f16", 2, ("tinyD", "tinyC"), "uniform", 702, 2),
    "alexnet_published": Config("alexnet_published", "bf16", 1, ("alexnet_published", "resnet18"), "normal", 703, 3),
}

ALL = dict(CONFIGS)
ALL.update(EXTRA)
ALL.update(PAPER_MIXES)
