"""MI355X-native slide step: ViT tile encoder + gated-attention MIL pool, forward and backward,
behind the C ABI of libslide.so (see include/slide.h; convolutional tile encoders: include/resnet.h).  This package is only the ctypes binding:
argument marshalling, nothing else.  There is no CPU fallback: importing `binding` without a
built libslide.so raises."""
from .binding import (SlideLib, SlideConfig, SlideError, config_from, lib_path,  # noqa: F401
                      ResNetLib, ResNetConfig, resnet_config_from)
