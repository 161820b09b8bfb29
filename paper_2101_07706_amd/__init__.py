"""MI355X-native skewed layer-wise neighbor sampling step for GCN training."""
