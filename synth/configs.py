"""The multi-tenant workloads and their seeded data.

Each configuration is a list of tenants that share one GPU.  Images are
224x224x3 tensors drawn from U[-1,1), standing in for the ImageNet-sized
inputs of the evaluation (Section 5.1, "Task and Benchmark"); no dataset is
read.  ``scale='small'`` swaps every tenant for a reduced member of the same
family (same operator kinds, ragged extents) for quick parity runs.
"""
from . import graphs as G

BASE_SEED = 20230411
TENANT_ID_STRIDE = 1 << 20
CONFIG_NAMES = {
    1: "toy-cnn(1)+toy-mlp(4) f32",
    2: "resnet18(8)+mobilenetv2(8) f32 224x224",
    3: "resnet50(16)+vgg16(8)+mobilenetv2(32) bf16 224x224",
    4: "2x{resnet18,resnet50,mobilenetv2,vgg16}(1) bf16 224x224",
    5: "bert-base-s128(8)+resnet50(32)+vgg16(16)+mobilenetv2(64) bf16",
    # a tenant mix of the evaluation itself (Section 5.2 and Table 2, "ALEX+V16+R18"; batch sizes are not stated there)
    6: "alexnet(8)+vgg16(8)+resnet18(8) f32 224x224",
    # "R50+V16+M3" and "R101+D121+M3" of the same table, the second one being the mix of more than 200 operators
    7: "resnet50(16)+vgg16(8)+mobilenetv3-large(32) bf16 224x224",
    8: "resnet101(8)+densenet121(8)+mobilenetv3-large(8) bf16 224x224",
}


def _tenants(config: int, scale: str):
    if config == 1:
        return [G.toy_cnn("f32", 1), G.toy_mlp("f32", 4)]
    if scale == "small":
        dt = "f32" if config == 2 else "bf16"
        if config == 2:
            return [G.small_resnet(dt, 3), G.small_mbv2(dt, 3)]
        if config == 3:
            return [G.small_resnet(dt, 4, bottleneck=True), G.small_cnn(dt, 3), G.small_mbv2(dt, 5)]
        if config == 4:
            return [G.small_resnet(dt, 1), G.small_resnet(dt, 1), G.small_resnet(dt, 1, bottleneck=True),
                    G.small_resnet(dt, 1, bottleneck=True), G.small_mbv2(dt, 1), G.small_mbv2(dt, 1),
                    G.small_cnn(dt, 1), G.small_cnn(dt, 1)]
        if config == 5:
            return [G.small_bert(dt, 3), G.small_resnet(dt, 4, bottleneck=True), G.small_cnn(dt, 2),
                    G.small_mbv2(dt, 6)]
        if config == 6:
            return [G.small_alexnet("f32", 3), G.small_cnn("f32", 2), G.small_resnet("f32", 3)]
        if config == 7:
            return [G.small_resnet(dt, 4, bottleneck=True), G.small_cnn(dt, 3), G.small_mbv3(dt, 5)]
        if config == 8:
            return [G.small_resnet(dt, 2, bottleneck=True), G.small_densenet(dt, 3), G.small_mbv3(dt, 2)]
    if config == 2:
        return [G.resnet18("f32", 8), G.mobilenetv2("f32", 8)]
    if config == 3:
        return [G.resnet50("bf16", 16), G.vgg16("bf16", 8), G.mobilenetv2("bf16", 32)]
    if config == 4:
        return [G.resnet18("bf16", 1), G.resnet18("bf16", 1), G.resnet50("bf16", 1), G.resnet50("bf16", 1),
                G.mobilenetv2("bf16", 1), G.mobilenetv2("bf16", 1), G.vgg16("bf16", 1), G.vgg16("bf16", 1)]
    if config == 5:
        return [G.bert_base("bf16", 8, 128), G.resnet50("bf16", 32), G.vgg16("bf16", 16),
                G.mobilenetv2("bf16", 64)]
    if config == 6:
        return [G.alexnet("f32", 8), G.vgg16("f32", 8), G.resnet18("f32", 8)]
    if config == 7:
        return [G.resnet50("bf16", 16), G.vgg16("bf16", 8), G.mobilenetv3_large("bf16", 32)]
    if config == 8:
        return [G.resnet101("bf16", 8), G.densenet121("bf16", 8), G.mobilenetv3_large("bf16", 8)]
    raise ValueError(f"unknown config {config}")


def build_config(config: int, scale: str = "full", with_data: bool = True):
    """Returns (tenants, data) where data[i] = (input, params) of tenant i,
    or (tenants, None) when ``with_data`` is false."""
    tenants = _tenants(config, scale)
    if not with_data:
        return tenants, None
    seed = BASE_SEED + (config - 1)
    data = [G.materialise(t, seed, i * TENANT_ID_STRIDE) for i, t in enumerate(tenants)]
    return tenants, data
