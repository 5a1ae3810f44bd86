"""MI355X-native RT-Lynx hot path: 2:4 activation-sparse linear layers (HIP, gfx950)."""
