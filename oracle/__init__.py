"""CPU oracle (test infrastructure): see vgg_ref.c and vgg_ref.py."""
