"""The benchmark configurations as plain dictionaries (shapes only; no arithmetic)."""

CONFIGS = {
    # tiny fp32 case the oracle finishes in seconds
    "tiny": dict(latent_channels=4, height=16, width=16, batch=1, channels=[32, 64], layers_per_block=1,
                 transformer_depth=[0, 0], mid_depth=1, head_dim=16, gn_groups=8, ctx_len=8, ctx_dim=32,
                 pooled_dim=0),
    # SD1.5/2.1-shaped UNet at 512px (latent 64x64), classifier-free guidance batch 2
    "sd_512": dict(latent_channels=4, height=64, width=64, batch=2, channels=[320, 640, 1280, 1280],
                   layers_per_block=2, transformer_depth=[1, 1, 1, 0], mid_depth=1, head_dim=64, gn_groups=32,
                   ctx_len=77, ctx_dim=1024, pooled_dim=0),
    # the metric configuration: same UNet at 768px (latent 96x96)
    "sd21_768": dict(latent_channels=4, height=96, width=96, batch=2, channels=[320, 640, 1280, 1280],
                     layers_per_block=2, transformer_depth=[1, 1, 1, 0], mid_depth=1, head_dim=64, gn_groups=32,
                     ctx_len=77, ctx_dim=1024, pooled_dim=0),
    # SDXL-shaped
    "sdxl_1024": dict(latent_channels=4, height=128, width=128, batch=2, channels=[320, 640, 1280],
                      layers_per_block=2, transformer_depth=[0, 2, 10], mid_depth=10, head_dim=64, gn_groups=32,
                      ctx_len=77, ctx_dim=2048, pooled_dim=1280),
    # reduced-width clone of the metric configuration (same topology, N=4 capable)
    "sd21_narrow": dict(latent_channels=4, height=24, width=24, batch=2, channels=[64, 128, 256, 256],
                        layers_per_block=2, transformer_depth=[1, 1, 1, 0], mid_depth=1, head_dim=64, gn_groups=32,
                        ctx_len=77, ctx_dim=1024, pooled_dim=0),
    # reduced-width clone of the SDXL-shaped model: no attention at level 0, deeper transformers below, pooled branch
    "sdxl_narrow": dict(latent_channels=4, height=32, width=32, batch=2, channels=[64, 128, 256],
                        layers_per_block=2, transformer_depth=[0, 1, 2], mid_depth=2, head_dim=64, gn_groups=32,
                        ctx_len=77, ctx_dim=256, pooled_dim=128),
    # video model: the 512px UNet over 16 frames (batch axis = frames, no guidance, one text embedding for all
    # frames) with a temporal attention layer (8 heads) after every spatial transformer
    "video_16f": dict(latent_channels=4, height=64, width=64, batch=16, channels=[320, 640, 1280, 1280],
                      layers_per_block=2, transformer_depth=[1, 1, 1, 0], mid_depth=1, head_dim=64, gn_groups=32,
                      ctx_len=77, ctx_dim=1024, pooled_dim=0, frames=16, temporal_heads=8),
    # reduced-width clone of the video model (same topology and frame count)
    "video_narrow": dict(latent_channels=4, height=16, width=16, batch=16, channels=[64, 128, 256, 256],
                         layers_per_block=2, transformer_depth=[1, 1, 1, 0], mid_depth=1, head_dim=64, gn_groups=32,
                         ctx_len=77, ctx_dim=1024, pooled_dim=0, frames=16, temporal_heads=8),
    # tiny video model for fp32 checks: 3 frames, attention at both levels
    "video_tiny": dict(latent_channels=4, height=8, width=8, batch=3, channels=[32, 64], layers_per_block=1,
                       transformer_depth=[1, 0], mid_depth=1, head_dim=16, gn_groups=8, ctx_len=8, ctx_dim=32,
                       pooled_dim=0, frames=3, temporal_heads=4),
}

RUNS = {
    "tiny": dict(N=2, T=10, w=1, S=1, sampler="ddim", cfg_scale=1.0, dtype="fp32"),
    "sd_512": dict(N=2, T=50, w=1, S=1, sampler="ddim", cfg_scale=7.5, dtype="bf16"),
    "sd21_768": dict(N=4, T=50, w=3, S=1, sampler="ddim", cfg_scale=7.5, dtype="bf16"),
    "sdxl_1024": dict(N=4, T=50, w=3, S=2, sampler="euler", cfg_scale=7.5, dtype="bf16"),
    "sd21_narrow": dict(N=4, T=50, w=3, S=1, sampler="ddim", cfg_scale=7.5, dtype="bf16"),
    "sdxl_narrow": dict(N=4, T=50, w=3, S=2, sampler="euler", cfg_scale=7.5, dtype="bf16"),
    "video_16f": dict(N=4, T=25, w=2, S=1, sampler="ddim", cfg_scale=1.0, dtype="bf16"),
    "video_narrow": dict(N=4, T=25, w=2, S=1, sampler="ddim", cfg_scale=1.0, dtype="bf16"),
    "video_tiny": dict(N=2, T=6, w=1, S=1, sampler="ddim", cfg_scale=1.0, dtype="fp32"),
}
