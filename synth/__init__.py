"""Seeded synthetic workloads (weights, inputs, arrival schedules).

Shared by the CPU oracle's tests and by the GPU library's binding; holds no
arithmetic of the forward pass."""
from .models import (ARCH_ENCODER, ARCH_MOBILENETV2, ARCH_NAMES, ARCH_RESNET50, ARCH_TINY_CNN, ARCH_VGG19, ARCH_VIT,
                     BN_EPS, ModelData, default_image_batch, encoder, image_batch, make_model,
                     mobilenet_v2, poisson_arrivals_ns, resnet50, tiny_cnn, token_batch, vgg19, vit)
from .container import pack

SEEDS = {ARCH_TINY_CNN: 0xC0FFEE + 1, ARCH_RESNET50: 0xC0FFEE + 2, ARCH_MOBILENETV2: 0xC0FFEE + 3,
         "colocation": 0xC0FFEE + 4, ARCH_ENCODER: 0xC0FFEE + 5, ARCH_VGG19: 0xC0FFEE + 6, ARCH_VIT: 0xC0FFEE + 7}
