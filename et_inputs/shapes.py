"""Encoder shapes of the synthetic workloads (a ViT in the SigLIP layout)."""
from dataclasses import dataclass, asdict


@dataclass(frozen=True)
class EncoderShape:
    n_layers: int
    d_model: int
    n_heads: int
    d_mlp: int
    patch: int
    image_h: int
    image_w: int
    channels: int = 3
    ln_eps: float = 1e-6
    has_final_ln: int = 1

    @property
    def grid_h(self):
        return self.image_h // self.patch

    @property
    def grid_w(self):
        return self.image_w // self.patch

    @property
    def tokens_per_frame(self):
        return self.grid_h * self.grid_w

    @property
    def head_dim(self):
        return self.d_model // self.n_heads

    @property
    def patch_dim(self):
        return self.channels * self.patch * self.patch

    def as_dict(self):
        return asdict(self)


# 4 layers, d=64, 4 heads of 16, MLP 256, 112x112 images -> 8x8 = 64 tokens per frame.
TINY = EncoderShape(n_layers=4, d_model=64, n_heads=4, d_mlp=256, patch=14,
                    image_h=112, image_w=112)

# SigLIP-so400m layout: 27 layers, d=1152, 16 heads of 72, MLP 4304, 384x384 -> 27x27 = 729.
SIGLIP = EncoderShape(n_layers=27, d_model=1152, n_heads=16, d_mlp=4304, patch=14,
                      image_h=384, image_w=384)
