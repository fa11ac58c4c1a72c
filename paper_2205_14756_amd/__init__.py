"""MI355X-native multi-scale linear attention (EfficientViT, Section 3.1)."""
