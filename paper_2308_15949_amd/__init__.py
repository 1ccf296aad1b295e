"""MI355X-native dynamic residual bottleneck (LAUDNet hot path): HIP kernels behind a C ABI
(include/laud.h, built into liblaud.so) and a thin ctypes binding.  Importing the package
does not load the library; the first call does, and raises if it has not been built."""
from . import inputs  # noqa: F401
from .binding import (  # noqa: F401
    BF16, F32, Bottleneck, Fmap, LaudError, abi_version, fmap_of, laud_channel_skip_conv,
    laud_dyn_bottleneck, laud_gather_patches, laud_layer_skip_compact, laud_mask_gen,
    laud_masker_dyn_bottleneck, laud_channel_masker, channel_masker_workspace,
    laud_dyn_bottleneck_unfused, dyn_bottleneck_unfused_workspace, laud_static_bottleneck,
    static_bottleneck_workspace, laud_stem, laud_stem3x3, stem_workspace, laud_dyn_projection_bottleneck,
    dyn_projection_workspace, GroupSE, laud_dyn_group_se_bottleneck, laud_dyn_group_se_projection_bottleneck, make_group_se,
    laud_stage_timing_enable, laud_stage_timing_read, load, laud_init, laud_dyn_bottleneck_noalloc, laud_probe_mfma, laud_probe_copy, laud_probe_read, laud_pack_weights, packed_weights_size,
    make_bottleneck, status_string, workspace_size,
)
