"""Seeded synthetic inputs and error measures shared by tests, smoke check and benchmark."""
