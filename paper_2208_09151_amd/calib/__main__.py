from . import build

print("built", build())
