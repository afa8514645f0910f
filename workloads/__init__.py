"""Seeded synthetic workloads shared by the CPU oracle's tests and the HIP path's tests.

This package holds network descriptions (the ORIGINAL strided patch CNNs) and
seeded random tensors only.  It contains none of the method's arithmetic: no
convolution, pooling, dilation planning, padding or loss code lives here.
"""
from .nets import Layer, Net, conv, maxpool, avgpool, CONFIGS, config_net  # noqa: F401
from .gen import (Workload, make_workload, make_params, pick_mask, sample_pixels,
                  config_workload)  # noqa: F401
from .video import (Layer3, VideoNet, VideoWorkload, VideoConfig, conv3, maxpool3, avgpool3,  # noqa: F401
                    make_video_workload, make_video_params, video_workload, VIDEO_CONFIGS,
                    TINY_VIDEO, STRIDED_VIDEO, CLIP_NET)
