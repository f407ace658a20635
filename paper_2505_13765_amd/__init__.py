"""MI355X-native WIND greedy decoder for RNN-T models: thin binding over libwind.so."""
from .binding import (WindError, WindModel, WindStats, lib_path, load_library)  # noqa: F401
