"""MI355X-native Big Little Decoder: HIP library (csrc/, built into libbild.so)
and its ctypes binding."""
from . import binding
from .binding import (ACCEPT_REJECTION, ACCEPT_THRESHOLD, BOTH, LARGE, SMALL, BildError, Model, ModelConfig, Pair, State, Stats,
                      config_from_shape, lib)
