"""MI355X-native masked-binary U-Net inference path (hand-written HIP for gfx950)."""
